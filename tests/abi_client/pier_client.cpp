// Plain client of the C ABI: no torch, no Python - hipMalloc'd buffers, raw pointers,
// hipStream_t handles.  Reads a case file written by the test, runs
//   H inner AdamW steps on each of G replicas -> resident outer step (Pier phase)
//   -> H more inner steps -> host-offload outer step (pinned anchor/M, three streams)
// and writes every buffer back for the test to compare with the oracle.
//
// case file (little endian): int32 n_tensors, G, H; int64 numel[n_tensors];
//   float theta0[N]; then for round in 0..1, step in 0..H-1, g in 0..G-1: float grad[N]
// result file: for g: theta_g[N], m_g[N], v_g[N]; anchor[N]; M[N]
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <vector>

#include "../../include/pier.h"

#define HIPCHECK(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) { fprintf(stderr, "%s: %s\n", #x, hipGetErrorString(e_)); return 2; } } while (0)
#define PIERCHECK(x) do { pier_status s_ = (x); if (s_ != PIER_OK) { fprintf(stderr, "%s: %s: %s\n", #x, pier_status_string(s_), pier_last_error()); return 3; } } while (0)

static bool read_all(FILE* f, void* p, size_t bytes) { return fread(p, 1, bytes, f) == bytes; }

int main(int argc, char** argv)
{
    if (argc != 3) { fprintf(stderr, "usage: pier_client <case file> <result file>\n"); return 1; }
    FILE* f = fopen(argv[1], "rb");
    if (!f) { perror("case file"); return 1; }
    int32_t hdr[3];
    if (!read_all(f, hdr, sizeof hdr)) return 1;
    const int nt = hdr[0], G = hdr[1], H = hdr[2];
    std::vector<int64_t> numel(nt);
    if (!read_all(f, numel.data(), sizeof(int64_t) * nt)) return 1;
    int64_t N = 0;
    for (int i = 0; i < nt; ++i) N += numel[i];
    std::vector<float> theta0(N), grad(N);
    if (!read_all(f, theta0.data(), sizeof(float) * N)) return 1;

    // one allocation per tensor and buffer kind, as a framework would hand them over
    auto alloc_list = [&](std::vector<float*>& v) -> int {
        v.assign(nt, nullptr);
        for (int i = 0; i < nt; ++i)
            if (numel[i] > 0) {
                HIPCHECK(hipMalloc(reinterpret_cast<void**>(&v[i]), sizeof(float) * numel[i]));
                HIPCHECK(hipMemset(v[i], 0, sizeof(float) * numel[i]));
            }
        return 0;
    };
    auto upload = [&](std::vector<float*>& v, const float* src) -> int {
        int64_t off = 0;
        for (int i = 0; i < nt; ++i) {
            if (numel[i] > 0) HIPCHECK(hipMemcpy(v[i], src + off, sizeof(float) * numel[i], hipMemcpyHostToDevice));
            off += numel[i];
        }
        return 0;
    };
    auto download = [&](std::vector<float*>& v, float* dst) -> int {
        int64_t off = 0;
        for (int i = 0; i < nt; ++i) {
            if (numel[i] > 0) HIPCHECK(hipMemcpy(dst + off, v[i], sizeof(float) * numel[i], hipMemcpyDeviceToHost));
            off += numel[i];
        }
        return 0;
    };

    std::vector<std::vector<float*>> P(G), M1(G), V(G), Gd(G);
    std::vector<float*> A, Mo;
    for (int g = 0; g < G; ++g) {
        if (alloc_list(P[g]) || alloc_list(M1[g]) || alloc_list(V[g]) || alloc_list(Gd[g])) return 2;
        if (upload(P[g], theta0.data())) return 2;
    }
    if (alloc_list(A) || alloc_list(Mo) || upload(A, theta0.data())) return 2;

    hipStream_t s_compute, s_in, s_out;
    HIPCHECK(hipStreamCreateWithFlags(&s_compute, hipStreamNonBlocking));
    HIPCHECK(hipStreamCreateWithFlags(&s_in, hipStreamNonBlocking));
    HIPCHECK(hipStreamCreateWithFlags(&s_out, hipStreamNonBlocking));

    pier_ctx* ctx = nullptr;
    PIERCHECK(pier_ctx_create(&ctx, nt, numel.data(), G));
    for (int g = 0; g < G; ++g)
        PIERCHECK(pier_bind_replica(ctx, g, P[g].data(), M1[g].data(), V[g].data(),
                                    reinterpret_cast<const void* const*>(Gd[g].data()), 0));
    PIERCHECK(pier_bind_outer(ctx, PIER_LOC_DEVICE, A.data(), Mo.data()));

    pier_adamw_hp hp = {3e-4f, 0.9f, 0.95f, 1e-8f, 0.1f, 1.0f, 0};
    pier_outer_hp ohp = {0.7f, 0.9f, PIER_PHASE_PIER};
    float *hA = nullptr, *hM = nullptr;
    void* workspace = nullptr;
    int64_t step = 0;
    for (int round = 0; round < 2; ++round) {
        for (int h = 0; h < H; ++h) {
            ++step;
            for (int g = 0; g < G; ++g) {
                if (!read_all(f, grad.data(), sizeof(float) * N)) return 1;
                HIPCHECK(hipStreamSynchronize(s_compute));   // the previous step still reads Gd[g]
                if (upload(Gd[g], grad.data())) return 2;
                hp.step = step;
                PIERCHECK(pier_inner_adamw(ctx, g, &hp, s_compute));
            }
        }
        if (round == 0) {
            PIERCHECK(pier_outer_step(ctx, &ohp, s_compute));
        } else {
            // move the outer state to pinned host memory and run the streamed step
            HIPCHECK(hipStreamSynchronize(s_compute));
            HIPCHECK(hipHostMalloc(reinterpret_cast<void**>(&hA), sizeof(float) * N, hipHostMallocDefault));
            HIPCHECK(hipHostMalloc(reinterpret_cast<void**>(&hM), sizeof(float) * N, hipHostMallocDefault));
            if (download(A, hA) || download(Mo, hM)) return 2;
            PIERCHECK(pier_bind_outer(ctx, PIER_LOC_HOST_PINNED, &hA, &hM));
            const size_t chunk = 4096;
            size_t wbytes = 0;
            PIERCHECK(pier_offload_workspace_bytes(ctx, chunk, &wbytes));
            HIPCHECK(hipMalloc(&workspace, wbytes));
            pier_offload_stats stats;
            ohp.outer_lr = 1.1f;
            PIERCHECK(pier_offload_stream(ctx, &ohp, chunk, workspace, wbytes, s_compute, s_in, s_out, &stats));
            fprintf(stderr, "offload: %d pieces, %d slots, %.3f ms\n", stats.n_pieces, stats.n_slots, stats.wall_ms);
        }
    }
    HIPCHECK(hipDeviceSynchronize());
    fclose(f);

    FILE* o = fopen(argv[2], "wb");
    if (!o) { perror("result file"); return 1; }
    std::vector<float> buf(N);
    for (int g = 0; g < G; ++g) {
        std::vector<float*>* lists[3] = {&P[g], &M1[g], &V[g]};
        for (auto* l : lists) {
            if (download(*l, buf.data())) return 2;
            fwrite(buf.data(), sizeof(float), N, o);
        }
    }
    fwrite(hA, sizeof(float), N, o);
    fwrite(hM, sizeof(float), N, o);
    fclose(o);
    PIERCHECK(pier_ctx_destroy(ctx));
    return 0;
}
