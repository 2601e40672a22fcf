// One speculative round through the C ABI alone (no Python, no PyTorch): reads a small problem
// from a binary file, runs k_max chained svip_draft_step calls and one svip_verify on buffers it
// allocates with hipMalloc, and prints the decisions as one JSON line.
//
// File layout (little endian): int32 B, k, V; float32 T, h; then float32 draft[B*k*V],
// target[B*(k+1)*V], u_sample[B*k], u_accept[B*k], u_resample[B].  V must be a multiple of 4.
#include <hip/hip_runtime.h>

#include <cstdio>
#include <cstdlib>
#include <vector>

#include "svip.h"

#define HIP_OK(x)                                                                   \
    do {                                                                            \
        hipError_t e_ = (x);                                                        \
        if (e_ != hipSuccess) {                                                     \
            std::fprintf(stderr, "%s: %s\n", #x, hipGetErrorString(e_));            \
            return 2;                                                               \
        }                                                                           \
    } while (0)
#define SVIP_OK_OR_DIE(x)                                                           \
    do {                                                                            \
        svip_status s_ = (x);                                                       \
        if (s_ != SVIP_OK) {                                                        \
            std::fprintf(stderr, "%s: %s\n", #x, svip_status_string(s_));           \
            return 3;                                                               \
        }                                                                           \
    } while (0)

template <typename T>
static bool read_vec(std::FILE *f, std::vector<T> &v, size_t n)
{
    v.resize(n);
    return std::fread(v.data(), sizeof(T), n, f) == n;
}

template <typename T>
static hipError_t to_device(const std::vector<T> &h, T **d)
{
    hipError_t e = hipMalloc(reinterpret_cast<void **>(d), h.size() * sizeof(T));
    if (e != hipSuccess) return e;
    return hipMemcpy(*d, h.data(), h.size() * sizeof(T), hipMemcpyHostToDevice);
}

int main(int argc, char **argv)
{
    if (argc != 2) {
        std::fprintf(stderr, "usage: %s problem.bin\n", argv[0]);
        return 1;
    }
    std::FILE *f = std::fopen(argv[1], "rb");
    if (!f) return 1;
    int hdr[3];
    float th[2];
    if (std::fread(hdr, sizeof(int), 3, f) != 3 || std::fread(th, sizeof(float), 2, f) != 2) return 1;
    const int B = hdr[0], k = hdr[1], V = hdr[2];
    const float T = th[0], h = th[1];
    if (B < 1 || k < 1 || V < 1 || V % 4 != 0) return 1;
    std::vector<float> draft, target, us, ua, ur;
    if (!read_vec(f, draft, (size_t)B * k * V) || !read_vec(f, target, (size_t)B * (k + 1) * V) ||
        !read_vec(f, us, (size_t)B * k) || !read_vec(f, ua, (size_t)B * k) || !read_vec(f, ur, (size_t)B))
        return 1;
    std::fclose(f);

    float *d_draft, *d_target, *d_us, *d_ua, *d_ur;
    HIP_OK(to_device(draft, &d_draft));
    HIP_OK(to_device(target, &d_target));
    HIP_OK(to_device(us, &d_us));
    HIP_OK(to_device(ua, &d_ua));
    HIP_OK(to_device(ur, &d_ur));
    int *d_tok, *d_len, *d_nacc, *d_next;
    double *d_lse;
    unsigned char *d_stop;
    void *ws;
    HIP_OK(hipMalloc(reinterpret_cast<void **>(&d_tok), sizeof(int) * B * k));
    HIP_OK(hipMalloc(reinterpret_cast<void **>(&d_lse), sizeof(double) * B * k));
    HIP_OK(hipMalloc(reinterpret_cast<void **>(&d_len), sizeof(int) * B));
    HIP_OK(hipMalloc(reinterpret_cast<void **>(&d_nacc), sizeof(int) * B));
    HIP_OK(hipMalloc(reinterpret_cast<void **>(&d_next), sizeof(int) * B));
    HIP_OK(hipMalloc(reinterpret_cast<void **>(&d_stop), B));
    HIP_OK(hipMemset(d_stop, 0, B));
    HIP_OK(hipMemset(d_tok, 0xFF, sizeof(int) * B * k));
    HIP_OK(hipMemset(d_len, 0, sizeof(int) * B));
    const size_t ws_bytes = svip_workspace_bytes(B, k, V);
    HIP_OK(hipMalloc(&ws, ws_bytes));
    hipStream_t st;
    HIP_OK(hipStreamCreate(&st));
    SVIP_OK_OR_DIE(svip_workspace_reset(ws, ws_bytes, st));

    // Algorithm 1's drafting loop: step j reads draft[:, j, :] and writes column j; flags stay on the device
    for (int j = 0; j < k; ++j)
        SVIP_OK_OR_DIE(svip_draft_step(d_draft + (size_t)j * V, SVIP_F32, B, V, (long long)k * V, T, h, j, k, d_us + j,
                                       d_stop, d_tok + j, nullptr, nullptr, d_lse + j, d_stop, d_len, k, ws, ws_bytes,
                                       st));
    SVIP_OK_OR_DIE(svip_verify(d_target, d_draft, SVIP_F32, B, k, V, (long long)(k + 1) * V, (long long)k * V, V, T, d_tok,
                               d_len, d_lse, d_ua, d_ur, d_nacc, d_next, nullptr, ws, ws_bytes, st));
    unsigned flags = 0;
    SVIP_OK_OR_DIE(svip_workspace_flags(ws, st, &flags));      // synchronises the stream

    std::vector<int> tok((size_t)B * k), len(B), nacc(B), next(B);
    HIP_OK(hipMemcpy(tok.data(), d_tok, sizeof(int) * B * k, hipMemcpyDeviceToHost));
    HIP_OK(hipMemcpy(len.data(), d_len, sizeof(int) * B, hipMemcpyDeviceToHost));
    HIP_OK(hipMemcpy(nacc.data(), d_nacc, sizeof(int) * B, hipMemcpyDeviceToHost));
    HIP_OK(hipMemcpy(next.data(), d_next, sizeof(int) * B, hipMemcpyDeviceToHost));
    std::printf("{\"flags\": %u, \"draft_len\": [", flags);
    for (int b = 0; b < B; ++b) std::printf("%s%d", b ? ", " : "", len[b]);
    std::printf("], \"n_accepted\": [");
    for (int b = 0; b < B; ++b) std::printf("%s%d", b ? ", " : "", nacc[b]);
    std::printf("], \"next_token\": [");
    for (int b = 0; b < B; ++b) std::printf("%s%d", b ? ", " : "", next[b]);
    std::printf("], \"tokens\": [");
    for (int i = 0; i < B * k; ++i) std::printf("%s%d", i ? ", " : "", tok[i]);
    std::printf("]}\n");
    return 0;
}
