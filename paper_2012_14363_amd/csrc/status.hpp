// Status codes used inside the library; values match the TP_* enum of the public header.
#pragma once

namespace tp {

enum Status : int {
    kSuccess = 0,
    kErrType = 1,
    kErrCount = 2,
    kErrArg = 3,
    kErrTruncate = 4,
    kErrBuffer = 5,
    kErrOther = 6,
    kErrRange = 7,
};

}  // namespace tp
