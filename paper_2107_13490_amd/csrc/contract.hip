// placeholder until the MFMA contractions land
#include "common.hpp"
#include "context.hpp"
extern "C" int adapt_fxp_gemm(adapt_ctx *, int, int, int, int, int, const void *, adapt_fmt, int, const void *, adapt_fmt, int, void *, int, adapt_epilogue) { return ADAPT_EUNSUPPORTED; }
extern "C" int adapt_conv_fwd(adapt_ctx *, adapt_conv_desc, const void *, adapt_fmt, const void *, adapt_fmt, void *, adapt_epilogue) { return ADAPT_EUNSUPPORTED; }
extern "C" int adapt_conv_dgrad(adapt_ctx *, adapt_conv_desc, const void *, adapt_fmt, const void *, adapt_fmt, void *, adapt_epilogue) { return ADAPT_EUNSUPPORTED; }
extern "C" int adapt_conv_wgrad(adapt_ctx *, adapt_conv_desc, const void *, adapt_fmt, const void *, adapt_fmt, void *, adapt_epilogue) { return ADAPT_EUNSUPPORTED; }
