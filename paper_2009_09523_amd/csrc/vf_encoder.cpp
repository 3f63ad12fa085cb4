// Placeholder until the encoder launch sequence lands.
#include "vf_ctx.h"
namespace vf {
std::unique_ptr<Model> make_encoder(const vf_config&) { return nullptr; }
}  // namespace vf
