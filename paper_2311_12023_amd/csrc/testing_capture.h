// State of lq_test_capture_iterate (testing build only): which configuration's iterate the next lq_error_table call of
// this host thread copies out.
#pragma once

namespace lq {
namespace testing {

struct Capture {
  bool armed = false;
  int cfg = -1;          // index into the call's configuration list
  int iter = 0;          // iteration whose quantized component is written out (dense)
  float* Q = nullptr;    // device, d x k
  double* sigma = nullptr;   // host, rank values: singular values of the Factorize that follows that iteration
};
Capture& capture();      // per host thread

}  // namespace testing
}  // namespace lq
