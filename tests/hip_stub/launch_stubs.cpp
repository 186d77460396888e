// No-op replacements for the kernel launchers: the sanitizer build exercises the host code around them.
#include "kvx_dev.h"
namespace kvx {
void launch_attention(const KvxBatch&, int, hipStream_t, hipEvent_t, hipEvent_t) {}
void launch_attention16(const KvxBatch&, hipStream_t, hipEvent_t, hipEvent_t) {}
void launch_combine(const KvxBatch&, hipStream_t) {}
void launch_pool(const KvxBatch&, hipStream_t) {}
void launch_score(const KvxBatch&, int, hipStream_t) {}
void launch_select(const KvxBatch&, int, hipStream_t) {}
void launch_rebuild_k(const KvxBatch&, int, hipStream_t) {}
void launch_rebuild_v(const KvxBatch&, int, hipStream_t) {}
void launch_append_bf16(const KvxBatch&, hipStream_t) {}
void launch_check_finite(const KvxBatch&, hipStream_t) {}
}  // namespace kvx
