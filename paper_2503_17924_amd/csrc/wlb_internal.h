// Internal declarations shared by the translation units of libwlb (not installed).
#pragma once
#include <cstdarg>
#include <cstddef>
#include <cstdint>

#include "wlb.h"

namespace wlb {

// Records the text returned by wlb_last_error() on this thread and passes `st` through.
wlb_status fail(wlb_status st, const char* fmt, ...);

constexpr int kGroupRows = 64;    // rows per schedule group (granularity of hull / full-range data)
constexpr int kFwdTileRows = 128; // query rows per forward / dQ work item
constexpr int kBwdKeyTile = 128;  // keys per dK/dV work item

inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

constexpr int kLists = 8;         // XCDs: workgroup b runs on XCD b % 8
#ifndef WLB_DKV_SPLIT
#define WLB_DKV_SPLIT 8
#endif
constexpr int kDkvSplit = WLB_DKV_SPLIT;      // a dK/dV item is at most 1/kDkvSplit of the mean load of a compute unit

// compute units of the GPU (256 when none is present: layout queries on the host)
int compute_units();
// bytes of the dK/dV partial results that follow delta / lse2 in the backward workspace
size_t dkv_partial_bytes(const wlb_attn_desc& d, const wlb_plan_layout& L);

// Validates desc; on success fills the plan layout.
wlb_status check_desc(const wlb_attn_desc* d);
void plan_layout(const wlb_attn_desc& d, wlb_plan_layout* L);

// Device-side launchers (defined in the .hip files); all asynchronous on `stream`.
wlb_status launch_plan(const wlb_attn_desc& d, const wlb_plan_layout& L, const int32_t* q_idx,
                       const int32_t* cu_seqlens_k, char* ws, void* stream);
wlb_status launch_fwd(const wlb_attn_desc& d, const wlb_plan_layout& L, const void* q, const void* k,
                      const void* v, void* o, float* lse, char* ws, void* stream);
wlb_status launch_bwd(const wlb_attn_desc& d, const wlb_plan_layout& L, const void* q, const void* k,
                      const void* v, const void* o, const float* lse, const void* d_o, void* dq,
                      void* dk, void* dv, char* ws, size_t off_delta, void* stream);

}  // namespace wlb
