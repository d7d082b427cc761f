// The gzip pass over the server's first message of a conversation (Sec. 4.2: that message carries the activations
// of the whole prompt, so it is compressed after quantisation).  Host-side byte work on a message that is on its
// way to the network anyway: DEFLATE in the gzip container (RFC 1951 / RFC 1952) through zlib, the system's
// implementation of that published format.  No device code in this file.
#include "../../include/moa.h"
#include "moa_common.h"

#include <limits.h>
#include <string.h>
#include <zlib.h>

extern "C" {

int32_t moa_msg_gzip_bound(size_t n, size_t *bytes_host)
{
    if (!bytes_host) return moa::api_fail(MOA_ERR_NULL, "msg_gzip_bound: bytes_host is NULL");
    if (n > (size_t)UINT_MAX / 2) return moa::api_fail(MOA_ERR_RANGE, "msg_gzip_bound: messages are limited to 2 GiB");
    // zlib's own worst case for one stream plus the 18 bytes of gzip header and trailer
    *bytes_host = (size_t)compressBound((uLong)n) + 18;
    return MOA_OK;
}

int32_t moa_msg_gzip(const void *msg_host, size_t n, void *out_host, size_t cap, size_t *out_bytes_host)
{
    if ((!msg_host && n) || !out_host || !out_bytes_host) return moa::api_fail(MOA_ERR_NULL, "msg_gzip: NULL pointer");
    if (n > (size_t)UINT_MAX / 2 || cap > (size_t)UINT_MAX) return moa::api_fail(MOA_ERR_RANGE, "msg_gzip: messages are limited to 2 GiB");
    z_stream zs;
    memset(&zs, 0, sizeof(zs));
    // window 15 + 16: the gzip container; header fields stay empty (no name, no time), so the bytes depend on the
    // message alone
    if (deflateInit2(&zs, Z_DEFAULT_COMPRESSION, Z_DEFLATED, 15 + 16, 8, Z_DEFAULT_STRATEGY) != Z_OK)
        return moa::api_fail(MOA_ERR_HIP, "msg_gzip: zlib would not start");
    static const unsigned char nothing = 0;
    zs.next_in = (Bytef *)(n ? msg_host : &nothing);
    zs.avail_in = (uInt)n;
    zs.next_out = (Bytef *)out_host;
    zs.avail_out = (uInt)cap;
    const int rc = deflate(&zs, Z_FINISH);
    const size_t produced = zs.total_out;
    deflateEnd(&zs);
    if (rc != Z_STREAM_END) return moa::api_fail(MOA_ERR_RANGE, "msg_gzip: output buffer too small (moa_msg_gzip_bound gives a size that always fits)");
    *out_bytes_host = produced;
    return MOA_OK;
}

int32_t moa_msg_gunzip(const void *gz_host, size_t n, void *out_host, size_t cap, size_t *out_bytes_host)
{
    if (!gz_host || (!out_host && cap) || !out_bytes_host) return moa::api_fail(MOA_ERR_NULL, "msg_gunzip: NULL pointer");
    if (n > (size_t)UINT_MAX || cap > (size_t)UINT_MAX) return moa::api_fail(MOA_ERR_RANGE, "msg_gunzip: messages are limited to 2 GiB");
    z_stream zs;
    memset(&zs, 0, sizeof(zs));
    if (inflateInit2(&zs, 15 + 16) != Z_OK) return moa::api_fail(MOA_ERR_HIP, "msg_gunzip: zlib would not start");
    unsigned char spare = 0;                   // an empty message still needs somewhere to point
    zs.next_in = (Bytef *)gz_host;
    zs.avail_in = (uInt)n;
    zs.next_out = (Bytef *)(cap ? out_host : &spare);
    zs.avail_out = (uInt)cap;
    const int rc = inflate(&zs, Z_FINISH);
    const size_t produced = zs.total_out;
    const bool out_full = zs.avail_out == 0, in_left = zs.avail_in > 0;
    inflateEnd(&zs);
    if (rc == Z_STREAM_END) {                  // the trailer's CRC-32 and length have been checked by zlib
        *out_bytes_host = produced;
        return MOA_OK;
    }
    // stopped before the end of the stream: out of output space with input still waiting, or out of input
    if ((rc == Z_BUF_ERROR || rc == Z_OK) && out_full && in_left)
        return moa::api_fail(MOA_ERR_RANGE, "msg_gunzip: output buffer too small for the message");
    return moa::api_fail(MOA_ERR_SHAPE, "msg_gunzip: not a complete, intact gzip stream");
}

}  // extern "C"
