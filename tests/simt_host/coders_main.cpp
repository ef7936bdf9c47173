// Runs the library's stream coders -- the real entry points of the sparse / predictive storage and of the
// Huffman stage, decoders and encoders, their kernels compiled for the CPU against the stand-in
// hip_runtime.h of this folder -- on cases read from a file, with every buffer
// allocated at exactly the size the call is told, so that AddressSanitizer sees any access the kernels'
// index arithmetic lets out of bounds.  TEST INFRASTRUCTURE ONLY (test_decoder_bounds_host.py).
//
// case file: uint32 count, then per case
//   'H' : uint64 n, stream_bytes, out_cap; stream bytes
//   'E' : uint64 n; the bytes to encode (result: the stream's bytes in use, then the two totals)
//   'Z' : int32 dtype, window; int64 maps, h, w; float tau, eps; the maps (result: info, uint64 totals[4], values and index bytes in use)
//   'S' : int32 dtype, window; int64 maps, h, w; float eps; uint64 info_bytes, values_bytes, indices_bytes; the three arrays
// result file: per case int32 status, uint64 out bytes, the output.
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

#include "../../include/fedhybrid.h"

namespace {

void* exact(size_t bytes)                                     // 16-byte aligned, sized to the byte (0 -> a 16-byte dummy)
{
    void* p = nullptr;
    if (posix_memalign(&p, 16, bytes ? bytes : 16) != 0) std::abort();
    std::memset(p, 0xA5, bytes ? bytes : 16);
    return p;
}

template <typename T> T take(FILE* f)
{
    T v;
    if (std::fread(&v, sizeof v, 1, f) != 1) { std::fprintf(stderr, "short case file\n"); std::exit(2); }
    return v;
}
void* take_bytes(FILE* f, size_t bytes)
{
    void* p = exact(bytes);
    if (bytes && std::fread(p, 1, bytes, f) != bytes) { std::fprintf(stderr, "short case file\n"); std::exit(2); }
    return p;
}
void put_result(FILE* f, int32_t status, const void* out, uint64_t bytes)
{
    std::fwrite(&status, sizeof status, 1, f);
    std::fwrite(&bytes, sizeof bytes, 1, f);
    if (bytes) std::fwrite(out, 1, bytes, f);
}

}  // namespace

int main(int argc, char** argv)
{
    if (argc != 3) { std::fprintf(stderr, "usage: %s cases results\n", argv[0]); return 2; }
    FILE* in = std::fopen(argv[1], "rb");
    FILE* out = std::fopen(argv[2], "wb");
    if (!in || !out) { std::fprintf(stderr, "cannot open files\n"); return 2; }
    const uint32_t count = take<uint32_t>(in);
    for (uint32_t c = 0; c < count; ++c) {
        const char kind = take<char>(in);
        if (kind == 'H') {
            const uint64_t n = take<uint64_t>(in), stream_bytes = take<uint64_t>(in), out_cap = take<uint64_t>(in);
            void* stream = take_bytes(in, stream_bytes);
            void* dst = exact(out_cap);
            const fh_status st = fh_huffman_decode(stream, stream_bytes, n, dst, out_cap, nullptr);
            put_result(out, (int32_t)st, dst, st == FH_OK ? out_cap : 0);
            std::free(stream);
            std::free(dst);
        } else if (kind == 'E') {
            const uint64_t n = take<uint64_t>(in);
            void* bytes = take_bytes(in, n);
            const size_t cap = fh_huffman_stream_bytes(n), ws_bytes = fh_huffman_workspace_bytes(n);
            void* stream = exact(cap);
            void* ws = exact(ws_bytes);
            uint64_t* totals = static_cast<uint64_t*>(exact(16));
            const fh_status st = fh_huffman_encode(bytes, n, stream, cap, totals, ws, ws_bytes, nullptr);
            std::vector<unsigned char> result;
            if (st == FH_OK) {
                result.assign(static_cast<unsigned char*>(stream), static_cast<unsigned char*>(stream) + totals[0]);
                result.insert(result.end(), reinterpret_cast<unsigned char*>(totals), reinterpret_cast<unsigned char*>(totals) + 16);
            }
            put_result(out, (int32_t)st, result.data(), result.size());
            std::free(bytes); std::free(stream); std::free(ws); std::free(totals);
        } else if (kind == 'Z') {
            const int32_t dtype = take<int32_t>(in), window = take<int32_t>(in);
            const int64_t maps = take<int64_t>(in), h = take<int64_t>(in), w = take<int64_t>(in);
            const float tau = take<float>(in), eps = take<float>(in);
            const size_t esize = dtype == FH_F32 ? 4u : 2u, numel = (size_t)(maps * h * w);
            void* x = take_bytes(in, numel * esize);
            const size_t info_bytes = fh_sparse_info_bytes(maps, h, w, window), index_cap = fh_sparse_index_bytes(maps, h, w, window);
            const size_t ws_bytes = fh_sparse_workspace_bytes(maps, h, w, window);
            void* info = exact(info_bytes);
            void* values = exact(numel * esize);
            void* indices = exact(index_cap);
            void* ws = exact(ws_bytes);
            uint64_t* totals = static_cast<uint64_t*>(exact(32));
            const fh_status st = fh_sparse_encode(x, (fh_dtype)dtype, maps, h, w, window, tau, eps, info, info_bytes, values,
                                                  numel * esize, indices, index_cap, totals, ws, ws_bytes, nullptr);
            std::vector<unsigned char> result;
            if (st == FH_OK) {
                const auto add = [&](const void* p, size_t n) { result.insert(result.end(), (const unsigned char*)p, (const unsigned char*)p + n); };
                add(info, info_bytes);
                add(totals, 32);
                add(values, (size_t)totals[0] * esize);
                add(indices, (size_t)totals[1]);
            }
            put_result(out, (int32_t)st, result.data(), result.size());
            std::free(x); std::free(info); std::free(values); std::free(indices); std::free(ws); std::free(totals);
        } else if (kind == 'S') {
            const int32_t dtype = take<int32_t>(in), window = take<int32_t>(in);
            const int64_t maps = take<int64_t>(in), h = take<int64_t>(in), w = take<int64_t>(in);
            const float eps = take<float>(in);
            const uint64_t info_bytes = take<uint64_t>(in), values_bytes = take<uint64_t>(in), indices_bytes = take<uint64_t>(in);
            void* info = take_bytes(in, info_bytes);
            void* values = take_bytes(in, values_bytes);
            void* indices = take_bytes(in, indices_bytes);
            const size_t out_bytes = (size_t)(maps * h * w) * (dtype == FH_F32 ? 4u : 2u);
            const size_t ws_bytes = fh_sparse_workspace_bytes(maps, h, w, window);
            void* dst = exact(out_bytes);
            void* ws = exact(ws_bytes);
            const fh_status st = fh_sparse_decode(info, values, values_bytes, indices, indices_bytes, (fh_dtype)dtype, maps, h, w,
                                                  window, eps, dst, out_bytes, ws, ws_bytes, nullptr);
            put_result(out, (int32_t)st, dst, st == FH_OK ? out_bytes : 0);
            std::free(info); std::free(values); std::free(indices); std::free(dst); std::free(ws);
        } else {
            std::fprintf(stderr, "unknown case kind\n");
            return 2;
        }
        std::fflush(out);
    }
    std::fclose(in);
    std::fclose(out);
    return 0;
}
