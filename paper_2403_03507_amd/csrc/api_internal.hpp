// Host-side helpers shared by the translation units of the C ABI (api.hip: context and step; api_stages.hip: the
// stateless stage calls; api_two_sided.hip: the two-sided rule of Definition 3.6): status / message plumbing and
// the argument checks every entry point runs before it launches anything.
#pragma once
#include "../../include/galore.h"
#include "common.hpp"

#include <cstddef>

struct galore_ctx;

namespace galore {
namespace api {

constexpr size_t kAlign = 256;
inline size_t align_up(size_t x) { return (x + kAlign - 1) / kAlign * kAlign; }

// Records the message (in ctx when given, and in the calling thread's slot read by galore_last_error(NULL)) and returns s.
galore_status fail(galore_ctx* ctx, galore_status s, const char* fmt, ...);
galore_status hip_fail(galore_ctx* ctx, hipError_t e, const char* where);
galore_status check_hparams(galore_ctx* ctx, const galore_hparams* hp);
galore_status check_matrix(galore_ctx* ctx, const galore_tensor& t, const char* what, int idx, bool need_data, bool allow_u8 = false);
galore_status check_weight_shape(galore_ctx* ctx, const galore_hparams& hp, const galore_tensor& w, int idx);

}  // namespace api
}  // namespace galore
