#include "model.h"
namespace speca {
Error make_dit_model(const speca_model_desc&, const speca_weights*, std::unique_ptr<Model>*) {
  SPECA_FAIL(SPECA_EUNSUPPORTED, "DiT model not built yet");
}
}
