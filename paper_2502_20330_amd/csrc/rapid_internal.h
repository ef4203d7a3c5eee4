// Internal declarations shared by the translation units of librapid.so.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "rapid.h"

struct rapid_ctx {
    int device;
    int n_cu;
    int last_hip_error;
    void* static_scratch;   // device address of this GPU's copy of the library's static scratch array
    int64_t accept_wait_ticks;   // bound of every inter-workgroup wait of the accept pass, 10 ns ticks
    int accept_slice;            // entries per workgroup of the accept row pass (0 = automatic)
    int probe_skew;              // streaming probe: 32nds of the mean share moved from odd to even workgroups
};

// ---- verify attention (verify_attn.hip)
struct AttnLaunch {
    const uint16_t* q;
    const uint16_t* k;
    const uint16_t* v;
    const int32_t* ctx_lens;
    const int32_t* gammas;
    const int32_t* page_table;
    uint16_t* out;
    float* lse_out;
    float* part_o;      // [B, Hkv, nsplit, RB*16, D] fp32, relative to part_m
    float* part_ml;     // [B, Hkv, nsplit, RB*16, 2] (running max in log2 units, sum)
    int32_t B, Qmax, Hq, Hkv, G, D, gamma;
    int32_t max_ctx;    // host bound of ctx_lens
    int32_t chunk, nsplit, RB;   // RB: 16-row blocks of the partials (wide: two teams of (RB + 1) / 2 and RB / 2 blocks)
    int32_t wide;       // 1: eight-wave kernel with two row teams
    int32_t rot;        // 1: dispatch slot x serves head (x + split) mod Hkv, 0: head x
    int32_t skew;       // tokens moved from the splits on odd dispatch slots to those on even ones
    int64_t bstride, tstride, hstride, pstride;   // elements
    int32_t page_shift, page_mask, max_pages;     // page_shift < 0: contiguous
    int32_t page_hi;    // largest page id the kernels will use (ids are clamped to [0, page_hi])
    float scale_log2e;
};
hipError_t launch_verify_attn(const AttnLaunch& a, hipStream_t stream);
hipError_t configure_verify_attn();   // per device, before the first launch
size_t attn_workspace_bytes(int B, int Hkv, int nsplit, int RB, int D);

// ---- accept pass (accept.hip)
struct AcceptLaunch {
    const float* zt;
    const float* zd;
    const int32_t* tokens;
    const int32_t* gammas;
    const float* uniforms;
    int32_t* n_accepted;
    int32_t* out_tokens;
    float* ratio;
    void* workspace;
    int32_t B, gmax, V;
    float eta, inv_T, tail_alpha;
    double inv_T_exact;   // 1 / (double)temperature
    // row statistics computed elsewhere (the output head's epilogue), or null:
    // (max z, sum exp((z - max)/T)) per chunk, [B*(gmax+1)][nch_t] and [B*gmax][nch_d] pairs
    const float* ext_t;
    const float* ext_d;
    int32_t nch_t, nch_d;
    int64_t wait_ticks;   // bound of an exchange wait in wall-clock ticks (100 MHz); 0 = never wait
    int32_t n_cu;         // compute units of the device (sizes the slices)
    int32_t force_nv;     // 2 / 4 / 8: slice of 4096 / 8192 / 16384 entries; 0 = automatic
};
hipError_t launch_accept(const AcceptLaunch& a, hipStream_t stream);
size_t accept_workspace_bytes(int B, int gmax, int V);
// the greedy limit T -> 0 (accept_greedy.hip); uses zt, zd, tokens, gammas, uniforms, outputs, workspace
hipError_t launch_accept_greedy(const AcceptLaunch& a, hipStream_t stream);
size_t accept_greedy_workspace_bytes(int B, int gmax, int V);

// ---- streaming-read probe (hbm_probe.hip)
hipError_t configure_hbm_read_probe();
hipError_t launch_hbm_read_probe(const rapid_ctx* ctx, const void* buf, size_t bytes, uint32_t* sink, hipStream_t stream);

// ---- output head (lm_head.hip)
struct LmHeadLaunch {
    const uint16_t* h;      // [n_rows][hidden] bf16
    const uint16_t* w;      // [vocab][hidden] bf16
    float* logits;          // [n_rows][ldz]
    float* stats;           // [n_rows][ceil(vocab / (16 nb))][2] or null
    int32_t n_rows, hidden, vocab;
    int32_t nb;             // 16-row vocabulary blocks per workgroup, 1..32 (statistics chunk = 16 nb)
    int64_t ldz;
    float inv_T;
};
hipError_t launch_lm_head(const LmHeadLaunch& a, hipStream_t stream);
hipError_t configure_lm_head();

// ---- cache bookkeeping (kv_cache.hip)
struct KvAppendLaunch {
    const uint16_t* k_new;      // [B][Qmax][Hkv][D]
    const uint16_t* v_new;
    const int32_t* ctx_lens;
    const int32_t* gammas;
    const int32_t* page_table;
    uint16_t* k_cache;
    uint16_t* v_cache;
    int32_t B, Qmax, Hkv, D, gamma;
    int32_t max_ctx;
    int64_t bstride, tstride, hstride, pstride;   // elements
    int32_t page_shift, page_mask, max_pages;     // page_shift < 0: contiguous
    int32_t page_hi;            // page ids are clamped to [0, page_hi]
};
struct KvCommitPagesLaunch {
    const int32_t* gammas;
    const int32_t* n_accepted;
    const int32_t* page_table;
    int32_t* ctx_lens;
    int32_t* released;          // [B][cap]
    int32_t* n_released;        // [B]
    int32_t B, Qmax, gamma, max_ctx, page_shift, max_pages, cap, page_hi;
};
hipError_t launch_kv_commit_pages(const KvCommitPagesLaunch& a, hipStream_t stream);
hipError_t launch_kv_append(const KvAppendLaunch& a, hipStream_t stream);
hipError_t launch_kv_commit(int B, int gamma, const int32_t* gammas, const int32_t* n_accepted, int32_t* ctx_lens,
                            hipStream_t stream);

// ---- retrieval chunk selection (retrieve.hip)
struct RetrieveLaunch {
    const float* emb;       // [n][dim]
    const float* query;     // [dim]
    float* sim;             // [n]
    int32_t* selected;      // [top_k], unused tail = -1
    int32_t* n_selected;    // [1]
    int32_t n, dim, top_k;
    float threshold;
};
hipError_t launch_retrieve(const RetrieveLaunch& a, hipStream_t stream);
