// Lloyd round for partition-scale k (k <= 64) and d in {64, 128}, fp32 embeddings: one kernel
// reads every embedding once, finds its nearest centroid and adds it to that centroid's sum.
//
// What it computes (EmbedPart paper, Alg. 3, step P <- KMeans(E, k)): the assignment
// argmin_j ||x - c_j||^2 = argmax_j (x.c_j - ||c_j||^2 / 2), lowest j on ties, and the per-cluster
// sums and counts from which the second pass forms the means.
//
// Mapping to the hardware (one wave = 64 lanes, lane = 16 * g + c):
//   * A wave owns a 16-point sub-tile.  Its rows are loaded from HBM with 16-byte loads that are
//     contiguous across the 16 lanes of a group (group g, step r reads point 4g + r), which is
//     also the operand layout of the update product.
//   * x.c runs on the fp32 matrix cores: v_mfma_f32_16x16x4_f32 with the points as the M
//     dimension and 16 centroids as the N dimension.  That operand needs lane c to hold point c,
//     so the sub-tile is transposed through a wave-private, padded LDS tile.
//   * The result holds, in lane (g, c), the scores of points 4g..4g+3 against centroid c; the
//     argmax is a 16-lane butterfly on (score, index).
//   * Sums: sums[centroid][column] += onehot[centroid][point] * x[point][column], again on the
//     matrix cores, contracted over the 16 points of the sub-tile.  Multiplying by exact 0/1
//     keeps every addition an ordinary fp32 addition in a fixed order; accumulators live in
//     registers for the whole life of the wave, so there are no atomics and no LDS traffic.
//   * At the end the four waves of a workgroup add their accumulators in wave order through LDS
//     and store one partial per workgroup; update_finalize_kernel reduces those in fp64.
#include <algorithm>

#include "kernels.h"

namespace ep {

namespace {

typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int kBlock = 256;
constexpr int kWaves = kBlock / 64;
constexpr int kSub = 16;  // points per sub-tile

enum Mode { kAssignOnly = 0, kUpdateOnly = 1, kFused = 2 };

__device__ __forceinline__ void wave_lds_fence() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

template <int D, int KT, int MODE>
__global__ __launch_bounds__(kBlock, (KT == 1 || (KT == 2 && D == 64)) ? 2 : 1) void lloyd_small_kernel(
    int64_t n, int64_t ld, int32_t k, int64_t subtiles_per_wg, const float *__restrict__ X,
    const float *__restrict__ C, const float *__restrict__ hneg, int32_t *__restrict__ labels_out,
    const int32_t *__restrict__ labels_in, float *__restrict__ min_d2, float *__restrict__ psum,
    int32_t *__restrict__ pcnt, double *__restrict__ obj_part) {
    constexpr int NJ = D / 16;       // 16-byte pieces per lane in the transposed layout; also column tiles
    constexpr int NH = D / 64;       // 16-byte pieces per lane and point in the load layout
    constexpr int STRIDE = D + 4;    // padded LDS row: consecutive rows start 4 banks apart
    __shared__ float lds[kWaves * kSub * STRIDE];
    __shared__ float xn_lds[kWaves][kSub];
    __shared__ double red[kWaves];
    __shared__ int32_t cnt_lds[16 * KT];

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int g = lane >> 4, c = lane & 15;
    float *tile = lds + wave * kSub * STRIDE;

    // Centroid operand of the assignment product: lane (g, c) holds, for centroid 16*mt + c,
    // columns 16j + 4g .. 16j + 4g + 3 for every j.  Padding centroids can never win.
    f32x4 creg[KT][NJ];
    float hn[KT];
    if (MODE != kUpdateOnly) {
#pragma unroll
        for (int mt = 0; mt < KT; ++mt) {
            const int cent = 16 * mt + c;
            const bool real = cent < k;
            hn[mt] = real ? hneg[cent] : -3.0e38f;
#pragma unroll
            for (int j = 0; j < NJ; ++j) {
                f32x4 v = {0.f, 0.f, 0.f, 0.f};
                if (real) v = *reinterpret_cast<const f32x4 *>(C + (int64_t)cent * D + 16 * j + 4 * g);
                creg[mt][j] = v;
            }
        }
    }

    f32x4 accu[KT][NJ];  // sums: lane (g, c), register v <-> centroid 16*mt + 4g + v, column col(t, c)
    int32_t cnt[KT];
#pragma unroll
    for (int mt = 0; mt < KT; ++mt) {
        cnt[mt] = 0;
#pragma unroll
        for (int t = 0; t < NJ; ++t) accu[mt][t] = f32x4{0.f, 0.f, 0.f, 0.f};
    }
    double obj_x = 0.0, obj_s = 0.0;

    const int64_t total_sub = (n + kSub - 1) / kSub;
    const int64_t first = (int64_t)blockIdx.x * subtiles_per_wg;
    const int64_t last = min(total_sub, first + subtiles_per_wg);

    f32x4 xcur[4][NH], xnext[4][NH];
    auto load_subtile = [&](int64_t st, f32x4(&dst)[4][NH]) {
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int64_t row = min(st * kSub + 4 * g + r, n - 1);  // rows past the end re-read the last row
#pragma unroll
            for (int h = 0; h < NH; ++h)
                dst[r][h] = *reinterpret_cast<const f32x4 *>(X + row * ld + 64 * h + 4 * c);
        }
    };

    int64_t st = first + wave;
    if (st < last) load_subtile(st, xcur);
    for (; st < last; st += kWaves) {
        const int64_t row0 = st * kSub;
        if (st + kWaves < last) load_subtile(st + kWaves, xnext);

        int32_t lab[4];
        if (MODE != kUpdateOnly) {
            // transpose through LDS: write point-major rows, read lane c <- point c
#pragma unroll
            for (int r = 0; r < 4; ++r)
#pragma unroll
                for (int h = 0; h < NH; ++h)
                    *reinterpret_cast<f32x4 *>(tile + (4 * g + r) * STRIDE + 64 * h + 4 * c) = xcur[r][h];
            wave_lds_fence();
            f32x4 areg[NJ];
#pragma unroll
            for (int j = 0; j < NJ; ++j) areg[j] = *reinterpret_cast<const f32x4 *>(tile + c * STRIDE + 16 * j + 4 * g);
            wave_lds_fence();  // the tile may be overwritten by the next sub-tile

            float xpart = 0.f;
#pragma unroll
            for (int j = 0; j < NJ; ++j)
                xpart += areg[j][0] * areg[j][0] + areg[j][1] * areg[j][1] + areg[j][2] * areg[j][2] +
                         areg[j][3] * areg[j][3];

            // scores: two accumulation chains per centroid tile (even / odd j), added at the end
            f32x4 acc0[KT], acc1[KT];
#pragma unroll
            for (int mt = 0; mt < KT; ++mt) {
                acc0[mt] = f32x4{hn[mt], hn[mt], hn[mt], hn[mt]};
                acc1[mt] = f32x4{0.f, 0.f, 0.f, 0.f};
            }
#pragma unroll
            for (int j = 0; j < NJ; j += 2)
#pragma unroll
                for (int e = 0; e < 4; ++e)
#pragma unroll
                    for (int mt = 0; mt < KT; ++mt) {
                        acc0[mt] = __builtin_amdgcn_mfma_f32_16x16x4f32(areg[j][e], creg[mt][j][e], acc0[mt], 0, 0, 0);
                        acc1[mt] = __builtin_amdgcn_mfma_f32_16x16x4f32(areg[j + 1][e], creg[mt][j + 1][e], acc1[mt],
                                                                         0, 0, 0);
                    }

            // argmax over centroids: inside the lane over tiles (ascending index), then over the row
            float bs[4];
            int32_t bi[4];
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                bs[v] = acc0[0][v] + acc1[0][v];
                bi[v] = c;
#pragma unroll
                for (int mt = 1; mt < KT; ++mt) {
                    const float s = acc0[mt][v] + acc1[mt][v];
                    if (s > bs[v]) { bs[v] = s; bi[v] = 16 * mt + c; }
                }
#pragma unroll
                for (int off = 8; off > 0; off >>= 1) {
                    const float os = __shfl_xor(bs[v], off, 64);
                    const int32_t oi = __shfl_xor(bi[v], off, 64);
                    if (os > bs[v] || (os == bs[v] && oi < bi[v])) { bs[v] = os; bi[v] = oi; }
                }
                lab[v] = (row0 + 4 * g + v < n) ? bi[v] : -1;
            }

            // lane c < 4 of every group owns point 4g + c for the stores and the objective
            const int sel = c & 3;
            const float my_s = sel == 0 ? bs[0] : sel == 1 ? bs[1] : sel == 2 ? bs[2] : bs[3];
            const int32_t my_l = sel == 0 ? lab[0] : sel == 1 ? lab[1] : sel == 2 ? lab[2] : lab[3];
            const int64_t my_row = row0 + 4 * g + c;
            const bool owner = c < 4 && my_row < n;
            if (owner) {
                labels_out[my_row] = my_l;
                obj_s += (double)my_s;
            }
            if (row0 + c < n) obj_x += (double)xpart;
            if (min_d2) {  // uniform branch
                float xn = xpart;
                xn += __shfl_xor(xn, 16, 64);
                xn += __shfl_xor(xn, 32, 64);
                if (g == 0) xn_lds[wave][c] = xn;
                wave_lds_fence();
                if (owner) min_d2[my_row] = fmaxf(xn_lds[wave][4 * g + c] - 2.f * my_s, 0.f);
                wave_lds_fence();
            }
        } else {
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int64_t row = row0 + 4 * g + v;
                const int32_t l = row < n ? labels_in[row] : -1;
                lab[v] = (l >= 0 && l < k) ? l : -1;
            }
        }

        if (MODE != kAssignOnly) {
#pragma unroll
            for (int r = 0; r < 4; ++r)
#pragma unroll
                for (int mt = 0; mt < KT; ++mt) {
                    const bool hit = lab[r] == 16 * mt + c;
                    const float a = hit ? 1.f : 0.f;
                    cnt[mt] += hit ? 1 : 0;
#pragma unroll
                    for (int t = 0; t < NJ; ++t)
                        accu[mt][t] = __builtin_amdgcn_mfma_f32_16x16x4f32(a, xcur[r][t >> 2][t & 3], accu[mt][t], 0, 0, 0);
                }
        }

#pragma unroll
        for (int r = 0; r < 4; ++r)
#pragma unroll
            for (int h = 0; h < NH; ++h) xcur[r][h] = xnext[r][h];
    }

    // ---- objective partial of this workgroup (fixed order) ----
    if (MODE != kUpdateOnly && obj_part) {
        double o = obj_x - 2.0 * obj_s;
        for (int off = 32; off > 0; off >>= 1) o += __shfl_down(o, off, 64);
        if (lane == 0) red[wave] = o;
    }

    // ---- partial sums of this workgroup: waves add their accumulators in wave order ----
    if (MODE != kAssignOnly) {
        __syncthreads();  // every wave has left its tile
        float *sums = lds;  // 16*KT x D floats
#pragma unroll 1
        for (int w = 0; w < kWaves; ++w) {
            if (wave == w) {
#pragma unroll
                for (int mt = 0; mt < KT; ++mt)
#pragma unroll
                    for (int t = 0; t < NJ; ++t)
#pragma unroll
                        for (int v = 0; v < 4; ++v) {
                            float *p = sums + (16 * mt + 4 * g + v) * D + 64 * (t >> 2) + 4 * c + (t & 3);
                            *p = (w == 0 ? 0.f : *p) + accu[mt][t][v];
                        }
            }
            __syncthreads();
        }
        for (int i = threadIdx.x; i < k * D; i += kBlock) psum[(int64_t)blockIdx.x * k * D + i] = sums[i];
        // counts: lanes of a column hold the counts of the 4 groups' points
        if (threadIdx.x < 16 * KT) cnt_lds[threadIdx.x] = 0;
        __syncthreads();
#pragma unroll
        for (int mt = 0; mt < KT; ++mt) {
            int32_t v = cnt[mt];
            v += __shfl_xor(v, 16, 64);
            v += __shfl_xor(v, 32, 64);
            if (g == 0 && v) atomicAdd(&cnt_lds[16 * mt + c], v);
        }
        __syncthreads();
        if ((int)threadIdx.x < k) pcnt[(int64_t)blockIdx.x * k + threadIdx.x] = cnt_lds[threadIdx.x];
    } else {
        __syncthreads();
    }
    if (MODE != kUpdateOnly && obj_part && threadIdx.x == 0) {
        double t = 0.0;
        for (int w = 0; w < kWaves; ++w) t += red[w];
        obj_part[blockIdx.x] = t;
    }
}

// hneg[j] = -||c_j||^2 / 2, accumulated in fp64.  One wave per centroid.
__global__ __launch_bounds__(kBlock) void half_norms_kernel(int32_t d, int32_t k, const float *__restrict__ C,
                                                             float *__restrict__ hneg) {
    const int j = blockIdx.x * kWaves + (threadIdx.x >> 6);
    if (j >= k) return;
    const int lane = threadIdx.x & 63;
    double acc = 0.0;
    for (int m = lane; m < d; m += 64) {
        const double v = (double)C[(int64_t)j * d + m];
        acc += v * v;
    }
    for (int off = 32; off > 0; off >>= 1) acc += __shfl_down(acc, off, 64);
    if (lane == 0) hneg[j] = (float)(-0.5 * acc);
}

// Second pass of a round.  Workgroup j forms centroid j: fp64 sum of the per-workgroup partials in
// workgroup order (two interleaved halves, added in a fixed order), divide, round to fp32; an
// empty cluster keeps its centroid.  It also leaves -||c_j||^2/2 for the next round and, in
// workgroup 0, the round's objective.
__global__ __launch_bounds__(kBlock) void lloyd_small_finalize_kernel(
    int32_t d, int32_t k, int parts, const float *__restrict__ psum, const int32_t *__restrict__ pcnt,
    const double *__restrict__ obj_part, int obj_parts, const float *__restrict__ C_prev, float *__restrict__ C_out,
    int64_t *__restrict__ counts, float *__restrict__ hneg, double *__restrict__ objective) {
    __shared__ double half_sum[kBlock];
    __shared__ float cn[128];
    __shared__ int64_t total_cnt;
    const int j = blockIdx.x, t = threadIdx.x;
    const int m = t % 128, half = t / 128;  // d <= 128
    if (t == 0) {
        int64_t cc = 0;
        for (int b = 0; b < parts; ++b) cc += pcnt[(int64_t)b * k + j];
        total_cnt = cc;
    }
    double s = 0.0;
    if (m < d)
        for (int b = half; b < parts; b += 2) s += (double)psum[((int64_t)b * k + j) * d + m];
    half_sum[t] = s;
    __syncthreads();
    if (half == 0 && m < d) {
        const double tot = half_sum[t] + half_sum[t + 128];
        const int64_t cc = total_cnt;
        const float cnew = cc > 0 ? (float)(tot / (double)cc) : C_prev[(int64_t)j * d + m];
        C_out[(int64_t)j * d + m] = cnew;
        cn[m] = cnew;
    }
    __syncthreads();
    if (t < 64) {  // same operations, in the same order, as half_norms_kernel
        double acc = 0.0;
        for (int mm = t; mm < d; mm += 64) {
            const double v = (double)cn[mm];
            acc += v * v;
        }
        for (int off = 32; off > 0; off >>= 1) acc += __shfl_down(acc, off, 64);
        if (t == 0) {
            hneg[j] = (float)(-0.5 * acc);
            counts[j] = total_cnt;
            if (j == 0 && objective) {
                double o = 0.0;
                for (int b = 0; b < obj_parts; ++b) o += obj_part[b];
                *objective = o;
            }
        }
    }
}

__global__ void sum_obj_kernel(const double *__restrict__ part, int count, double *__restrict__ out) {
    if (threadIdx.x == 0 && blockIdx.x == 0) {
        double t = 0.0;
        for (int b = 0; b < count; ++b) t += part[b];
        *out = t;
    }
}

struct Geometry {
    int blocks;
    int64_t subtiles_per_wg;
};

Geometry geometry(int64_t n) {
    const int64_t total_sub = ceil_div(n, kSub);
    int64_t wgs = std::min<int64_t>(kSmallMaxBlocks, ceil_div(total_sub, kWaves));
    const int64_t per = ceil_div(total_sub, wgs);
    return Geometry{(int)ceil_div(total_sub, per), per};
}

template <int MODE>
int launch_mode(const ep_problem &p, const float *X, const float *C, const KmeansWs &w, int32_t *labels_out,
                const int32_t *labels_in, float *min_d2, bool want_obj, hipStream_t s) {
    const Geometry geo = geometry(p.n);
    const int kt = p.k <= 16 ? 1 : p.k <= 32 ? 2 : 4;
    double *obj = want_obj ? w.obj_part : nullptr;
    ProfScope prof(MODE == kUpdateOnly ? EP_PROF_UPDATE_SUMS : EP_PROF_LLOYD_MAIN, s);
#define EP_SMALL_LAUNCH(D_, KT_)                                                                                   \
    lloyd_small_kernel<D_, KT_, MODE><<<geo.blocks, kBlock, 0, s>>>(p.n, p.ld, p.k, geo.subtiles_per_wg, X, C, w.cnorm, \
                                                                    labels_out, labels_in, min_d2, w.psum, w.pcnt, obj)
    if (p.d == 128) {
        if (kt == 1) EP_SMALL_LAUNCH(128, 1); else if (kt == 2) EP_SMALL_LAUNCH(128, 2); else EP_SMALL_LAUNCH(128, 4);
    } else {
        if (kt == 1) EP_SMALL_LAUNCH(64, 1); else if (kt == 2) EP_SMALL_LAUNCH(64, 2); else EP_SMALL_LAUNCH(64, 4);
    }
#undef EP_SMALL_LAUNCH
    EP_LAUNCH_CHECK();
    return EP_OK;
}

}  // namespace

bool small_path_supported(const ep_problem &p) {
    return p.dtype == EP_F32 && (p.d == 64 || p.d == 128) && p.k <= 64;
}

int small_blocks(const ep_problem &p) { return geometry(p.n).blocks; }

int launch_small_half_norms(const ep_problem &p, const float *C, const KmeansWs &w, hipStream_t s) {
    half_norms_kernel<<<(unsigned)ceil_div(p.k, kWaves), kBlock, 0, s>>>(p.d, p.k, C, w.cnorm);
    EP_LAUNCH_CHECK();
    return EP_OK;
}

int launch_small_assign(const ep_problem &p, const void *X, const float *C, const KmeansWs &w, int32_t *labels,
                        float *min_d2, double *objective, hipStream_t s) {
    int rc = launch_mode<kAssignOnly>(p, static_cast<const float *>(X), C, w, labels, nullptr, min_d2,
                                      objective != nullptr, s);
    if (rc != EP_OK) return rc;
    if (objective) {
        sum_obj_kernel<<<1, 64, 0, s>>>(w.obj_part, small_blocks(p), objective);
        EP_LAUNCH_CHECK();
    }
    return EP_OK;
}

int launch_small_finalize(const ep_problem &p, const float *C_prev, float *C_out, int64_t *counts,
                          const KmeansWs &w, double *objective, hipStream_t s) {
    const int parts = small_blocks(p);
    lloyd_small_finalize_kernel<<<p.k, kBlock, 0, s>>>(p.d, p.k, parts, w.psum, w.pcnt, w.obj_part, parts, C_prev,
                                                       C_out, counts, w.cnorm, objective);
    EP_LAUNCH_CHECK();
    return EP_OK;
}

int launch_small_update(const ep_problem &p, const void *X, const int32_t *labels, const float *C_prev,
                        float *C_out, int64_t *counts, const KmeansWs &w, hipStream_t s) {
    int rc = launch_mode<kUpdateOnly>(p, static_cast<const float *>(X), nullptr, w, nullptr, labels, nullptr, false, s);
    if (rc != EP_OK) return rc;
    return launch_small_finalize(p, C_prev, C_out, counts, w, nullptr, s);
}

int launch_small_round(const ep_problem &p, const void *X, float *C, const KmeansWs &w, int32_t *labels,
                       int64_t *counts, double *objective, hipStream_t s) {
    int rc = launch_mode<kFused>(p, static_cast<const float *>(X), C, w, labels, nullptr, nullptr,
                                 objective != nullptr, s);
    if (rc != EP_OK) return rc;
    return launch_small_finalize(p, C, C, counts, w, objective, s);
}

}  // namespace ep
