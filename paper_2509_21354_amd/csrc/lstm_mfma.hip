#include "common.hpp"
#include "kernels.hpp"
namespace kvev {
hipError_t launch_lstm_mfma(const LstmArgs &, hipStream_t) { return hipErrorNotSupported; }
}
