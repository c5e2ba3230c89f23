// Physical eviction (sections 3.2-3.3 of the paper: a chunk that is not kept is
// discarded, which is where the memory ratio n / (W + M) of section 3.3 comes
// from).  Per sequence a compact store holds at most k summaries, ascending by
// chunk id, with their ids and scores.  Freshly scored chunks (ids above every
// id in the store) are merged in and the best min(k, count + n_new) under the
// order of the top-k selection (score descending, NaN as minus infinity, ties to
// the lower id) stay.  A chunk that drops out can never return, because the
// scores of old chunks do not change, so the store always equals the top-k over
// every chunk seen so far.
//
// One workgroup per sequence.  Candidates are already in ascending id order
// (store entries, then the new chunks), so after ranking by counting, a kept
// candidate's new slot is the number of kept candidates before it: surviving
// store rows only move towards slot 0 and the new rows are appended.  Rows move
// in batches of destination slots: every source of a batch is read into
// registers before the batch is written, and a batch only overwrites slots
// below the sources that later batches still need.
#include "common.hpp"
#include "kernels.hpp"

namespace kvev {

typedef uint32_t piece_t __attribute__((ext_vector_type(4)));    // a 16-byte piece of a row

constexpr int kRetainBatch = 32;      // destination rows per pass (32 rows x up to 512 B = 16 B per thread x 4)

__global__ __launch_bounds__(256) void retain_kernel(RetainArgs a)
{
    extern __shared__ unsigned char smem_r[];
    const int s = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int cnt = min(max(a.count[s], 0), a.k_cap);
    const int n = cnt + a.n_new;
    float *s_key = reinterpret_cast<float *>(smem_r);                  // [n] ranking key
    float *s_raw = s_key + n;                                          // [n] score as stored (a NaN stays a NaN)
    int *s_src = reinterpret_cast<int *>(s_raw + n);                   // [k_cap] candidate that lands in each slot
    __shared__ int s_cnt[4];

    int32_t *ids = a.ids + (size_t)s * a.k_cap;
    float *uc = a.uc + (size_t)s * a.k_cap;
    const float *un = a.un + (size_t)s * a.n_new_cap;
    for (int c = tid; c < n; c += 256) {
        const float u = c < cnt ? uc[c] : un[c - cnt];
        s_raw[c] = u;
        s_key[c] = u != u ? -INFINITY : u;
    }
    __syncthreads();

    // rank by counting; the candidate index is the id order
    int base = 0;
    for (int c0 = 0; c0 < n; c0 += 256) {
        const int c = c0 + tid;
        bool keep = false;
        if (c < n) {
            const float u = s_key[c];
            int rank = 0;
            for (int j = 0; j < n; ++j) {
                const float uj = s_key[j];
                rank += (uj > u || (uj == u && j < c)) ? 1 : 0;
            }
            keep = rank < a.k;
        }
        const unsigned long long mask = __ballot(keep);
        if (lane == 0) s_cnt[wave] = __popcll(mask);
        __syncthreads();
        int before = base;
        for (int w = 0; w < wave; ++w) before += s_cnt[w];
        if (c < n) {
            const int pos = before + __popcll(mask & ((1ull << lane) - 1ull));
            if (keep) s_src[pos] = c;
        }
        base += s_cnt[0] + s_cnt[1] + s_cnt[2] + s_cnt[3];
        __syncthreads();
    }
    const int kept = base;             // <= k <= k_cap

    // ids and scores of the new store: through registers, then a barrier, then the write
    for (int p0 = 0; p0 < kept; p0 += 256) {
        const int p = p0 + tid;
        int id = 0;
        float u = 0.f;
        if (p < kept) {
            const int c = s_src[p];
            id = c < cnt ? ids[c] : a.first_chunk + (c - cnt);
            u = s_raw[c];
        }
        __syncthreads();               // slots [p0, p0+256) are sources only of slots >= p0: all read before any is written
        if (p < kept) { ids[p] = id; uc[p] = u; }
    }

    // rows: 16-byte pieces, kRetainBatch destination slots per pass
    const int vec_per_row = a.row_bytes / 16;
    unsigned char *Kc = static_cast<unsigned char *>(a.Kc) + (size_t)s * a.k_cap * a.row_bytes;
    unsigned char *Vc = static_cast<unsigned char *>(a.Vc) + (size_t)s * a.k_cap * a.row_bytes;
    const unsigned char *Kn = static_cast<const unsigned char *>(a.Kn) + (size_t)s * a.n_new_cap * a.row_bytes;
    const unsigned char *Vn = static_cast<const unsigned char *>(a.Vn) + (size_t)s * a.n_new_cap * a.row_bytes;
    constexpr int PIECES = kRetainBatch * 32 / 256;       // pieces per thread per tensor at 32 vectors per row
    for (int p0 = 0; p0 < kept; p0 += kRetainBatch) {
        piece_t rk[PIECES], rv[PIECES];
        const int pieces = min(kRetainBatch, kept - p0) * vec_per_row;
#pragma unroll
        for (int i = 0; i < PIECES; ++i) {
            const int e = tid + 256 * i;
            if (e < pieces) {
                const int p = p0 + e / vec_per_row, v = e % vec_per_row;
                const int c = s_src[p];
                const unsigned char *sk = c < cnt ? Kc + (size_t)c * a.row_bytes : Kn + (size_t)(c - cnt) * a.row_bytes;
                const unsigned char *sv = c < cnt ? Vc + (size_t)c * a.row_bytes : Vn + (size_t)(c - cnt) * a.row_bytes;
                rk[i] = *reinterpret_cast<const piece_t *>(sk + v * 16);
                rv[i] = *reinterpret_cast<const piece_t *>(sv + v * 16);
            }
        }
        __syncthreads();
#pragma unroll
        for (int i = 0; i < PIECES; ++i) {
            const int e = tid + 256 * i;
            if (e < pieces) {
                const int p = p0 + e / vec_per_row, v = e % vec_per_row;
                *reinterpret_cast<piece_t *>(Kc + (size_t)p * a.row_bytes + v * 16) = rk[i];
                *reinterpret_cast<piece_t *>(Vc + (size_t)p * a.row_bytes + v * 16) = rv[i];
            }
        }
        __syncthreads();
    }
    if (tid == 0) a.count[s] = kept;
}

hipError_t launch_retain(const RetainArgs &a, hipStream_t st)
{
    if (a.S == 0) return hipSuccess;
    const size_t n_max = (size_t)a.k_cap + a.n_new;
    const size_t lds = n_max * 2 * sizeof(float) + (size_t)a.k_cap * sizeof(int) + 16;
    hipLaunchKernelGGL(retain_kernel, dim3(a.S), dim3(256), lds, st, a);
    return hipGetLastError();
}

}  // namespace kvev
