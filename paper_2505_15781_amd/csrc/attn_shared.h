// Attention kernel for larger active sets: the NW (4 or 8) wavefronts of a workgroup share each K/V tile.
// Included by attention.hip (uses its helpers); head_dim 128 only.
//
// Work item = (sequence, kv head, block of NW*NQ query tiles of 16 rows, key slice). The workgroup
// streams its key slice in tiles of 64 keys: every thread fetches part of the K rows and of the V rows
// as they are stored (transposing LDS reads form the V operand of the second product), two LDS stages alternate, and the global
// loads of the next tile (with 8 wavefronts: of the next two) are in flight while the current one is multiplied. Each wavefront multiplies its own NQ query
// tiles against the shared tile, so a K or V fragment read from LDS feeds NQ MFMAs and the tile is read
// from L2 once per 64*NQ query rows instead of once per 16.
#pragma once

template <int NQ, int NW, bool ONCE>
__global__ __launch_bounds__(64 * NW, 8 / NW) __attribute__((amdgpu_waves_per_eu(2, 2))) void attn_bf16_shared(
    const bf16_t *__restrict__ Q, const bf16_t *__restrict__ Kc, const bf16_t *__restrict__ Vc,
    const int *__restrict__ row_off, bf16_t *__restrict__ out, float *__restrict__ part, int batch,
    int Hq, int Hkv, int L, int q_blocks, int splits, int tiles_per_split, int rows_cap,
    float scale_log2e) {
    constexpr int DH = 128, KT2 = 64;
    constexpr int K_STRIDE = DH * 2 + 16;      // bytes per key row
    constexpr int V_STRIDE = DH * 2 + 32;      // bytes per V row
    constexpr int K_BYTES = KT2 * K_STRIDE, STAGE_BYTES = K_BYTES + KT2 * V_STRIDE;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int G = Hq / Hkv;
    int pair, within;
    if (!attn_item(blockIdx.x, batch * Hkv, q_blocks * splits, pair, within)) return;
    const int split = within % splits, qb = within / splits;
    const int kvh = pair % Hkv, b = pair / Hkv;

    const int r0 = row_off[b], nrows = row_off[b + 1] - r0;
    const int nq = nrows * G;
    const int mb0 = qb * NW * NQ * 16;
    if (mb0 >= nq) return;                       // uniform for the workgroup

    const int qi = lane & 15, g = lane >> 4;
    bool q_ok[NQ];
    int q_row[NQ], q_head[NQ];
    bf16x8 qf[NQ][DH / 32];
#pragma unroll
    for (int j = 0; j < NQ; ++j) {
        const int mq = mb0 + (wave * NQ + j) * 16 + qi;
        q_ok[j] = mq < nq && r0 + mq / G < rows_cap;
        q_row[j] = q_ok[j] ? r0 + mq / G : 0;
        q_head[j] = kvh * G + (q_ok[j] ? mq % G : 0);
        const bf16_t *qp = Q + ((size_t)q_row[j] * Hq + q_head[j]) * DH + 8 * g;
#pragma unroll
        for (int ks = 0; ks < DH / 32; ++ks) {
            uint4 v = q_ok[j] ? *reinterpret_cast<const uint4 *>(qp + 32 * ks) : make_uint4(0, 0, 0, 0);
            qf[j][ks] = *reinterpret_cast<bf16x8 *>(&v);
        }
    }

    const bf16_t *Kb = Kc + ((size_t)b * Hkv + kvh) * (size_t)L * DH;
    const bf16_t *Vb = Vc + ((size_t)b * Hkv + kvh) * (size_t)L * DH;
    const int n_tiles = (L + KT2 - 1) / KT2;
    const int t0 = split * tiles_per_split, t1 = min(n_tiles, t0 + tiles_per_split);

    // per thread: CH chunks (16 B) of K and of V per tile, in register set A or B on their way to LDS
    constexpr int NT = 64 * NW, CH = KT2 * (DH / 8) / NT;
    uint4 kA[CH], vA[CH], kB[CH], vB[CH];
    // ONCE: one block of query tiles per (sequence, kv head), so nobody else reads these K/V rows in this launch and
    // they are fetched with the non-temporal hint; with several blocks they are meant to be found in L2 again.
    // The loads are unconditional (keys past the end are clamped to the last row: their scores are masked and their
    // probabilities are zero) so that the code is one straight line and the waits below can count: with a branch
    // around every load the compiler can only wait for all of them, which puts the loads of the tile after next in
    // front of the products they are meant to overlap.
    auto load_tile = [&](int t, uint4 (&kr)[CH], uint4 (&vr)[CH]) {
        const int key0 = t * KT2;
#pragma unroll
        for (int i = 0; i < CH; ++i) {
            const int c = tid + NT * i, key = c >> 4, ch = c & 15, gk = min(key0 + key, L - 1);
            if (ONCE) {
                kr[i] = load16_nt(Kb + (size_t)gk * DH + ch * 8);
                vr[i] = load16_nt(Vb + (size_t)gk * DH + ch * 8);
            } else {
                kr[i] = load16(Kb + (size_t)gk * DH + ch * 8);
                vr[i] = load16(Vb + (size_t)gk * DH + ch * 8);
            }
        }
    };
    auto store_tile = [&](int stage, const uint4 (&kr)[CH], const uint4 (&vr)[CH]) {
        unsigned char *ksm = smem_raw + stage * STAGE_BYTES, *vsm = ksm + K_BYTES;
#pragma unroll
        for (int i = 0; i < CH; ++i) {
            const int c = tid + NT * i, key = c >> 4, ch = c & 15;
            *reinterpret_cast<uint4 *>(ksm + key * K_STRIDE + ch * 16) = kr[i];
            *reinterpret_cast<uint4 *>(vsm + key * V_STRIDE + ch * 16) = vr[i];
        }
    };
    const int v_lane_off = (4 * g + (qi >> 2)) * V_STRIDE + (qi & 3) * 8;

    float m_run[NQ];
    f32x4 acc[NQ][DH / 16], l_acc[NQ];
    const bf16x8 ones = row_sum_operand(lane);
#pragma unroll
    for (int j = 0; j < NQ; ++j) {
        m_run[j] = -INFINITY;
        l_acc[j] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int i = 0; i < DH / 16; ++i) acc[j][i] = f32x4{0.f, 0.f, 0.f, 0.f};
    }

    // products and softmax of tile t, which sits in LDS stage `stage`
    auto multiply = [&](int t, int stage) {
        const unsigned char *ksm = smem_raw + stage * STAGE_BYTES, *vsm = ksm + K_BYTES;
        f32x4 st[NQ][4];
#pragma unroll
        for (int j = 0; j < NQ; ++j)
#pragma unroll
            for (int jt = 0; jt < 4; ++jt) st[j][jt] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int jt = 0; jt < 4; ++jt) {
            const unsigned char *krow = ksm + (16 * jt + qi) * K_STRIDE + g * 16;
#pragma unroll
            for (int ks = 0; ks < DH / 32; ++ks) {
                const bf16x8 kf = *reinterpret_cast<const bf16x8 *>(krow + ks * 64);
#pragma unroll
                for (int j = 0; j < NQ; ++j)
                    st[j][jt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf, qf[j][ks], st[j][jt], 0, 0, 0);
            }
        }
        // st[j][jt][i] is the score of key 16 jt + 4g + i of this tile against query qi of tile j
        bf16x8 pb[NQ][2];
#pragma unroll
        for (int j = 0; j < NQ; ++j)
            softmax_step<4, DH / 16>(st[j], m_run[j], l_acc[j], acc[j], pb[j], t * KT2 + 4 * g, L, (t + 1) * KT2 > L,
                                     scale_log2e);
#pragma unroll
        for (int hh = 0; hh < 2; ++hh)
#pragma unroll
            for (int j = 0; j < NQ; ++j)
                l_acc[j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ones, pb[j][hh], l_acc[j], 0, 0, 0);
#pragma unroll
        for (int hh = 0; hh < 2; ++hh)
#pragma unroll
            for (int mt = 0; mt < DH / 16; ++mt) {
                const bf16x8 av = vt_operand(vsm + v_lane_off, mt, V_STRIDE, 32 * hh);
#pragma unroll
                for (int j = 0; j < NQ; ++j)
                    acc[j][mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av, pb[j][hh], acc[j][mt], 0, 0, 0);
            }
    };

    // Tile t0 + i is multiplied out of LDS stage i & 1. t0 and t1 are uniform for the workgroup, so every
    // wavefront passes the same barriers. The steady-state loops issue the same loads on every pass, without a
    // branch around them, so the wait in front of a tile store counts exactly that tile's loads (behind a
    // conditional load the compiler can only wait for everything, which would put the prefetch in front of the
    // products it is meant to overlap); the last tiles, which prefetch less, are peeled off.
    if (t0 < t1) {
        load_tile(t0, kA, vA);
        store_tile(0, kA, vA);
        int t = t0;
        if (NW == 8) {
            // one workgroup per compute unit: while a tile is multiplied, the next one waits in one register set
            // and the one after it is being fetched into the other (16 registers per set)
            if (t + 1 < t1) load_tile(t + 1, kA, vA);
            __syncthreads();
            for (; t + 3 < t1; t += 2) {
                load_tile(t + 2, kB, vB);
                multiply(t, 0);
                store_tile(1, kA, vA);
                __syncthreads();
                load_tile(t + 3, kA, vA);
                multiply(t + 1, 1);
                store_tile(0, kB, vB);
                __syncthreads();
            }
            // one to three tiles are left: t in stage 0, t + 1 on its way in set A
            if (t + 2 < t1) load_tile(t + 2, kB, vB);
            multiply(t, 0);
            if (t + 1 < t1) {
                store_tile(1, kA, vA);
                __syncthreads();
                multiply(t + 1, 1);
                if (t + 2 < t1) {
                    store_tile(0, kB, vB);
                    __syncthreads();
                    multiply(t + 2, 0);
                }
            }
        } else {
            // two workgroups per compute unit cover each other's waits: one tile ahead is enough
            __syncthreads();
            for (; t + 1 < t1; ++t) {
                const int stage = (t - t0) & 1;
                load_tile(t + 1, kA, vA);
                multiply(t, stage);
                store_tile(stage ^ 1, kA, vA);
                __syncthreads();
            }
            multiply(t, (t - t0) & 1);
        }
    }

#pragma unroll
    for (int j = 0; j < NQ; ++j) {
        const float l = query_lanes_sum(l_acc[j][0]);
        if (!q_ok[j]) continue;
        if (splits == 1) {
            const float inv = 1.f / l;
            bf16_t *op = out + ((size_t)q_row[j] * Hq + q_head[j]) * DH;
#pragma unroll
            for (int mt = 0; mt < DH / 16; ++mt) {
                uint2 w;
                w.x = (uint32_t)f2bf(acc[j][mt][0] * inv) | ((uint32_t)f2bf(acc[j][mt][1] * inv) << 16);
                w.y = (uint32_t)f2bf(acc[j][mt][2] * inv) | ((uint32_t)f2bf(acc[j][mt][3] * inv) << 16);
                *reinterpret_cast<uint2 *>(op + 16 * mt + 4 * g) = w;
            }
        } else {
            float *rec = part + (((size_t)q_row[j] * Hq + q_head[j]) * splits + split) * (DH + 4);
            if (g == 0) {
                rec[0] = m_run[j];
                rec[1] = l;
            }
#pragma unroll
            for (int mt = 0; mt < DH / 16; ++mt) *reinterpret_cast<f32x4 *>(rec + 4 + 16 * mt + 4 * g) = acc[j][mt];
        }
    }
}
