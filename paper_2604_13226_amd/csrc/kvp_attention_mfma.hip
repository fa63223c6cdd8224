// placeholder until the MFMA kernel lands
#include "kvp_device.h"
namespace kvp {
int launch_attention_mfma(const AttnArgs &, void *) { return (int)hipErrorNotSupported; }
}
